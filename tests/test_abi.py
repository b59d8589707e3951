"""The C-ABI library loads without a GPU and exports every function include/swarm.h declares.
Host-side argument validation is exercised where it needs no device."""
import ctypes
import os
import re

import pytest

from paper_2603_17803_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "swarm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swarm_[a-z_]+)\s*\(", text)))


def test_header_and_binding_agree_on_the_export_list():
    assert declared_functions() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    lib = binding.load()
    for name in declared_functions():
        assert hasattr(lib, name), name
        assert ctypes.cast(getattr(lib, name), ctypes.c_void_p).value


def test_library_was_built_from_the_sources_on_disk():
    """The library is git-ignored but travels with the tree: its compiled-in source hash must be the hash of
    csrc/ and include/swarm.h as they are now, or the GPU tests would exercise an older binary."""
    binding.load()
    assert binding.library_is_current(), "libswarm.so is older than its sources: run __graft_entry__.build()"


def test_null_context_is_rejected_without_touching_a_device():
    lib = binding.load()
    assert lib.swarm_destroy(None) == binding.SWARM_EINVAL
    assert binding.swarm_score_select(0, 0, 0, 1, 1, 8, 1, 0, 1, 1, 0, None) == binding.SWARM_EINVAL
    assert binding.swarm_coact_accumulate(0, 0, 1, 1, 1, 1, 0, 65536, 0) == binding.SWARM_EINVAL
    assert binding.swarm_map_requests(0, 0, 1, 1, 1, 1, 0, 1, 0, 1, 1, None, None, 0, 0, 0, 1) == binding.SWARM_EINVAL


def test_struct_layout_matches_the_header():
    # kind(4) pad(4) data(8) H N d G (4 each) = 32 bytes on LP64
    assert ctypes.sizeof(binding.swarm_keys) == 32
    assert binding.swarm_keys.data.offset == 8 and binding.swarm_keys.H.offset == 16


def test_create_fails_cleanly_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(binding.SwarmError):
        binding.swarm_create(0, 0)
    with pytest.raises(RuntimeError):
        binding.Swarm(0)
