"""The Python layer checks what the C ABI cannot see -- dtype, size, layout and device of every
tensor -- and raises before the call.  CPU only: a rejected call never reaches the library's kernels
(the wrong-dtype and short-buffer cases are reported before the device is looked at, so CPU
tensors serve)."""
import pytest
import torch

from paper_1407_4764_amd import binding


def _f(*shape):
    return torch.zeros(shape, dtype=torch.float32)


def _ws(n=1 << 22):
    return torch.zeros(n, dtype=torch.uint8)


def test_int64_row_numbers_are_rejected():
    """torch.randint gives int64; read as int32 pairs half the batch would silently become row 0."""
    w, Xp, Xn = _f(16), _f(8, 16), _f(8, 16)
    i64 = torch.zeros(4, dtype=torch.int64)
    i32 = torch.zeros(4, dtype=torch.int32)
    with pytest.raises(TypeError, match="idx_pos"):
        binding.svm_sgd_step(w, None, Xp, i64, Xn, i32, 1.0, 1, False, _ws())
    with pytest.raises(TypeError, match="idx_neg"):
        binding.svm_sgd_step(w, None, Xp, i32, Xn, i64, 1.0, 1, False, _ws())
    with pytest.raises(TypeError, match="idx_pos"):
        binding.svm_sgd_pass(w, None, Xp, i64.reshape(2, 2), Xn, i32.reshape(2, 2), 1.0, 1, False, _ws())
    with pytest.raises(ValueError, match="columns"):
        binding.svm_sgd_step(w, None, _f(8, 12), i32, Xn, i32, 1.0, 1, False, _ws())


def test_short_or_mistyped_ranking_buffers_are_rejected():
    X, w = _f(1000, 16), _f(16)
    with pytest.raises(ValueError, match="all_scores"):
        binding.rank_dense(X, w, None, 10, _ws(), all_scores=_f(999))
    with pytest.raises(TypeError, match="all_scores"):
        binding.rank_dense(X, w, None, 10, _ws(), all_scores=torch.zeros(1000, dtype=torch.float64))
    with pytest.raises(ValueError, match="ws"):
        binding.rank_dense(X, w, None, 10, _ws(1024))
    with pytest.raises(ValueError, match="out scores"):
        binding.rank_dense(X, w, None, 10, _ws(), out=(_f(1, 5), torch.zeros((1, 10), dtype=torch.int32)))
    with pytest.raises(TypeError, match="out indices"):
        binding.rank_dense(X, w, None, 10, _ws(), out=(_f(1, 10), torch.zeros((1, 10), dtype=torch.int64)))
    with pytest.raises(TypeError, match="X"):
        binding.rank_dense(X.double(), w, None, 10, _ws())
    with pytest.raises(ValueError, match="W"):
        binding.rank_dense(X, _f(12), None, 10, _ws())
    with pytest.raises(ValueError, match="bias"):
        binding.rank_dense(X, _f(3, 16), _f(2), 10, _ws())
    with pytest.raises(ValueError, match="out scores"):
        binding.rank_dense_noalloc(X, w, None, 10, (_f(1, 5), torch.zeros((1, 10), dtype=torch.int32)))


def test_code_stores_must_have_their_own_dtypes():
    with pytest.raises(TypeError, match="codes"):
        binding.rank_pq(torch.zeros((100, 16), dtype=torch.int32), _f(16, 256), 0.0, 5, _ws())
    with pytest.raises(ValueError, match="lut"):
        binding.rank_pq(torch.zeros((100, 16), dtype=torch.uint8), _f(8, 256), 0.0, 5, _ws())
    with pytest.raises(TypeError, match="bits"):
        binding.rank_binary(torch.zeros((100, 4), dtype=torch.int64), 128, _f(128), 0.0, 5, _ws())
    with pytest.raises(ValueError, match="bits"):
        binding.rank_binary(torch.zeros((100, 4), dtype=torch.int32), 256, _f(256), 0.0, 5, _ws())
    with pytest.raises(ValueError, match="w holds"):
        binding.rank_binary(torch.zeros((100, 4), dtype=torch.int32), 128, _f(64), 0.0, 5, _ws())
    with pytest.raises(TypeError, match="scores"):
        binding.topk(torch.zeros(100, dtype=torch.float16), 5, _ws())
    with pytest.raises(TypeError, match="codes"):
        binding.pq_encode(_f(10, 32), _f(4, 256, 8), _ws(), codes=torch.zeros((10, 4), dtype=torch.int32))


def test_host_tensors_are_rejected_when_everything_else_is_right():
    with pytest.raises(ValueError, match="GPU memory"):
        binding.rank_dense(_f(1000, 16), _f(16), None, 10, _ws())
    with pytest.raises(ValueError, match="GPU memory"):
        binding.topk(_f(1000), 10, _ws())
