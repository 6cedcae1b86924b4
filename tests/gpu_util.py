"""GPU-side helpers for the parity tests: move a case to the device in the
K x M / N x M layout, call the C ABI, bring C back as M x N."""
import numpy as np


def _torch():
    import torch
    return torch


def to_dev_KM(A16, lda=None):
    """A (M x K fp16) -> device tensor K x lda holding A^T; padding is NaN."""
    torch = _torch()
    M, K = A16.shape
    lda = lda or (M + 7) // 8 * 8
    At = np.full((K, lda), np.nan, np.float16)
    At[:, :M] = A16.T
    return torch.from_numpy(At).cuda(), lda


def new_C(N, M, ldc=None, fill=float("nan")):
    torch = _torch()
    ldc = ldc or (M + 7) // 8 * 8
    return torch.full((N, ldc), fill, dtype=torch.float16, device="cuda"), ldc


def run_tw(tw, packed, A16, N, *, lda=None, ldc=None, fill=float("nan")):
    """Returns (C as M x N float64, raw N x ldc fp16 array)."""
    torch = _torch()
    M = A16.shape[0]
    At, lda = to_dev_KM(A16, lda)
    Ct, ldc = new_C(N, M, ldc, fill)
    tw.tw_gemm(At.data_ptr(), M, lda, tw.LAYOUT_KM, packed, Ct.data_ptr(), ldc,
               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Ct.cpu().numpy()
    return raw[:, :M].T.astype(np.float64), raw


def run_dense(tw, A16, B16, *, lda=None, ldb=None, ldc=None):
    torch = _torch()
    M, K = A16.shape
    N = B16.shape[1]
    At, lda = to_dev_KM(A16, lda)
    ldb = ldb or (N + 7) // 8 * 8
    Bp = np.full((K, ldb), np.nan, np.float16)
    Bp[:, :N] = B16
    Bd = torch.from_numpy(Bp).cuda()
    Ct, ldc = new_C(N, M, ldc)
    tw.tw_dense_gemm(At.data_ptr(), Bd.data_ptr(), Ct.data_ptr(), M, K, N, lda, ldb, ldc,
                     tw.LAYOUT_KM, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Ct.cpu().numpy()
    return raw[:, :M].T.astype(np.float64), raw


def run_tw_mk(tw, packed, A16, N, *, lda=None, ldc=None, fill=float("nan")):
    """Row-major layout: A is M x lda, C is M x ldc."""
    torch = _torch()
    M, K = A16.shape
    lda = lda or (K + 7) // 8 * 8
    ldc = ldc or (N + 7) // 8 * 8
    Ap = np.full((M, lda), np.nan, np.float16)
    Ap[:, :K] = A16
    Ad = torch.from_numpy(Ap).cuda()
    Cd = torch.full((M, ldc), fill, dtype=torch.float16, device="cuda")
    tw.tw_gemm(Ad.data_ptr(), M, lda, tw.LAYOUT_MK, packed, Cd.data_ptr(), ldc,
               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Cd.cpu().numpy()
    return raw[:, :N].astype(np.float64), raw


def run_dense_mk(tw, A16, B16):
    torch = _torch()
    M, K = A16.shape
    N = B16.shape[1]
    lda, ldb, ldc = (K + 7) // 8 * 8, (N + 7) // 8 * 8, (N + 7) // 8 * 8
    Ap = np.zeros((M, lda), np.float16); Ap[:, :K] = A16
    Bp = np.zeros((K, ldb), np.float16); Bp[:, :N] = B16
    Ad, Bd = torch.from_numpy(Ap).cuda(), torch.from_numpy(Bp).cuda()
    Cd = torch.full((M, ldc), float("nan"), dtype=torch.float16, device="cuda")
    tw.tw_dense_gemm(Ad.data_ptr(), Bd.data_ptr(), Cd.data_ptr(), M, K, N, lda, ldb, ldc,
                     tw.LAYOUT_MK, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return Cd.cpu().numpy()[:, :N].astype(np.float64)


PAD8 = 0x55      # padding byte of int8 operands: any use of it shows up in the sums


def to_dev_KM_i8(A8, lda=None):
    """A (M x K int8) -> device tensor K x lda holding A^T."""
    torch = _torch()
    M, K = A8.shape
    lda = lda or (M + 15) // 16 * 16
    At = np.full((K, lda), PAD8, np.int8)
    At[:, :M] = A8.T
    return torch.from_numpy(At).cuda(), lda


def new_C_i8(N, M, c_dtype, ldc=None, fill=-77):
    torch = _torch()
    ldc = ldc or (M + 15) // 16 * 16
    dt = torch.int8 if c_dtype else torch.int32
    return torch.full((N, ldc), fill, dtype=dt, device="cuda"), ldc


def run_tw_i8(tw, packed, A8, N, *, c_dtype=0, scale=1.0, lda=None, ldc=None, fill=-77):
    """Returns (C as M x N int64, raw N x ldc array)."""
    torch = _torch()
    M = A8.shape[0]
    At, lda = to_dev_KM_i8(A8, lda)
    Ct, ldc = new_C_i8(N, M, c_dtype, ldc, fill)
    tw.tw_gemm_i8(At.data_ptr(), M, lda, packed, Ct.data_ptr(), ldc, c_dtype, scale,
                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Ct.cpu().numpy()
    return raw[:, :M].T.astype(np.int64), raw


def run_dense_i8(tw, A8, B8, *, c_dtype=0, scale=1.0, lda=None, ldb=None, ldc=None, fill=-77):
    torch = _torch()
    M, K = A8.shape
    N = B8.shape[1]
    At, lda = to_dev_KM_i8(A8, lda)
    ldb = ldb or (N + 15) // 16 * 16
    Bp = np.full((K, ldb), PAD8, np.int8)
    Bp[:, :N] = B8
    Bd = torch.from_numpy(Bp).cuda()
    Ct, ldc = new_C_i8(N, M, c_dtype, ldc, fill)
    tw.tw_dense_gemm_i8(At.data_ptr(), Bd.data_ptr(), Ct.data_ptr(), M, K, N, lda, ldb, ldc, c_dtype, scale,
                        torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    raw = Ct.cpu().numpy()
    return raw[:, :M].T.astype(np.int64), raw


def run_conv(tw, packed, X16, geom, N, *, ldc=None, fill=float("nan")):
    """Implicit-img2col launch: X16 is C x ldx (wide layout).  Returns (C over the wide grid as
    Mp x N float64, raw N x ldc fp16 array)."""
    torch = _torch()
    Mp = geom.Mp
    Xd = torch.from_numpy(np.ascontiguousarray(X16)).cuda()
    b = tw.tw_conv_bind(packed, geom, X16.shape[1])
    Ct, ldc = new_C(N, Mp, ldc, fill)
    tw.tw_conv_gemm(Xd.data_ptr(), b, Ct.data_ptr(), ldc, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    b.free()
    raw = Ct.cpu().numpy()
    return raw[:, :Mp].T.astype(np.float64), raw


def run_conv_i8(tw, packed, X8, geom, N, *, c_dtype=0, scale=1.0, ldc=None, fill=-77):
    """Implicit-img2col launch on int8: X8 is C x ldx (wide layout).  Returns (C over the wide grid
    as Mp x N int64, raw N x ldc array)."""
    torch = _torch()
    Mp = geom.Mp
    Xd = torch.from_numpy(np.ascontiguousarray(X8)).cuda()
    b = tw.tw_conv_bind(packed, geom, X8.shape[1])
    Ct, ldc = new_C_i8(N, Mp, c_dtype, ldc, fill)
    tw.tw_conv_gemm_i8(Xd.data_ptr(), b, Ct.data_ptr(), ldc, c_dtype, scale, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    b.free()
    raw = Ct.cpu().numpy()
    return raw[:, :Mp].T.astype(np.int64), raw
