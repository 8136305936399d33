"""The C ABI used from C++ with nothing but include/hac.h and the HIP runtime."""
import ctypes as C
import os

import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hac():
    import paper_2108_12704_amd as lib
    lib.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    return lib


def test_c_abi_client_without_python_or_torch(hac):
    """tests/native/abi_client.cpp: a C++ client of include/hac.h that allocates with hipMalloc and
    checks hac_dot, shac_dot and hac_forward against host loops; here only its entry point is called."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "libabi_client.so")
    assert os.path.exists(path), "tests/native/libabi_client.so is not built (python __graft_entry__.py builds it)"
    torch.cuda.synchronize()
    client = C.CDLL(path)
    client.abi_client_run.argtypes = [C.c_char_p, C.c_size_t]
    msg = C.create_string_buffer(256)
    rc = client.abi_client_run(msg, 256)
    assert rc == 0, f"step {rc}: {msg.value.decode()}"
