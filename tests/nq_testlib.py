"""Shared plumbing of the GPU parity tests: run the same seeded inputs through the HIP path
(via the C ABI binding) and through the CPU oracle.  No arithmetic of the method lives here: the
quantised test inputs below are the seeded float draws of the input module put through the oracle's
quantiser (Eq. 1)."""
import numpy as np
import torch

from oracle import nq_oracle as oracle
from paper_2506_17870_amd import inputs


def weights(N, K, sigma, n_bits=8, seed=0):
    """INT-n codes [N,K] of N(0, sigma) weights and their per-output-channel steps fp32[N] (oracle, Eq. 1)."""
    return oracle.quantize(inputs.float_weights(N, K, sigma, seed), n_bits)


def tensor_codes(a, n_bits=8):
    """Per-tensor quantisation of an activation tensor (oracle, Eq. 1 with the whole tensor as one row)."""
    codes, step = oracle.quantize(np.ascontiguousarray(a, np.float32).reshape(1, -1), n_bits)
    return codes.reshape(a.shape), np.float32(step[0])


def relu_activations(shape, seed=0):
    return tensor_codes(inputs.relu_floats(shape, seed))


def gaussian_activations(shape, seed=0):
    return tensor_codes(inputs.gaussian_floats(shape, seed))


def plan_weights(ops, n_bits=8, seed=0):
    """(codes, steps, bias) of every conv / fc of a network plan: the plan's float weights through the oracle."""
    from paper_2506_17870_amd import network
    return [None if w is None else oracle.quantize(w[0], n_bits) + (w[1],)
            for w in network.plan_float_weights(ops, seed)]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


class Case:
    """One nested layer: int8 weights [N,K] + scales, prepared on both sides."""

    def __init__(self, nq, w_int, scale, n_bits, l_bits):
        self.nq, self.n, self.l = nq, n_bits, l_bits
        self.w_int, self.scale = w_int, scale
        self.N, self.K = w_int.shape
        self.cfg = nq.make_cfg(n_bits, l_bits)
        self.W = nq.NestedWeight.from_int8(dev(w_int), dev(scale), self.cfg)
        # oracle side, from its own pages
        self.o_high, self.o_low = oracle.decompose_pack(w_int, n_bits, l_bits)
        self.ow_full = oracle.weights_from_pages(self.o_high, self.o_low, self.N, self.K, n_bits, l_bits)
        self.ow_part = oracle.weights_from_pages(self.o_high, None, self.N, self.K, n_bits, l_bits)

    def pages_match(self):
        return (np.array_equal(host(self.W.high)[:self.o_high.size], self.o_high) and
                np.array_equal(host(self.W.low)[:self.o_low.size], self.o_low))


# Kernel choices every case is run with: the library's own, then each kernel forced through nq_set_tuning
# (1 generic, 2 windowed, 3 register-stationary, 4 large GEMM, 5 few input channels, 6 few rows, 9 stationary
# weights; a kernel
# that does not apply to a shape is not forced, the library's choice runs again).  The large-GEMM kernel is
# also run with every tile height it is built for (rows per block = 32 * TM, TM = 2..5): the library picks
# the height from the shape, so without this a parity shape reaches one height only ("tm6": 128 rows with the
# compute unit to itself; "tm7": 128 rows x 128 columns per block).
KERNEL_CHOICES = ("", "1", "2", "3", "4", "4/tm2", "4/tm3", "4/tm4", "4/tm5", "4/tm6", "4/tm7", "5", "6", "9")


def set_choice(choice):
    import paper_2506_17870_amd as nq
    kernel, _, tm = choice.partition("/tm")
    nq.nq_set_tuning(nq.NQ_TUNE_KERNEL, int(kernel) if kernel else 0)
    nq.nq_set_tuning(nq.NQ_TUNE_BIG_TM, int(tm) if tm else 0)


def each_kernel(choices=KERNEL_CHOICES):
    for k in choices:
        set_choice(k)
        try:
            yield k
        finally:
            set_choice("")


def epi_pair(nq, case, full, M_shape, s_a=1.0, bias=None, residual=None, s_r=0.0, relu=False, out_int8=False,
             inv_s_out=1.0, dump=True):
    """Builds the device epilogue descriptor + holders, and the oracle kwargs.  dump=False leaves the
    accumulator dump out, which is what lets the library pick its vector epilogues."""
    N = case.N
    keep = {}
    keep["acc"] = torch.empty(tuple(M_shape) + (N,), dtype=torch.int32, device="cuda") if dump else None
    keep["bias"] = dev(bias) if bias is not None else None
    keep["res"] = dev(residual) if residual is not None else None
    epi = nq.make_epilogue(s_a, keep["bias"], keep["res"], s_r, relu, out_int8, inv_s_out, keep["acc"])
    okw = dict(s_a=s_a, s_w=case.scale, part_l_bits=0 if full else case.l, bias=bias, residual=residual,
               s_r=s_r, relu=relu, out_int8=out_int8, inv_s_out=inv_s_out)
    return epi, keep, okw


def check_outputs(y_gpu, acc_gpu, y_ref, acc_ref, out_int8):
    if acc_gpu is not None:
        assert np.array_equal(acc_gpu, acc_ref), "int32 accumulators differ"
    if out_int8:
        assert np.array_equal(y_gpu, y_ref), "requantised int8 outputs differ"
    else:
        # tolerance of the fp32 outputs: 1e-5 relative (they are in fact expected to be identical)
        denom = np.maximum(np.abs(y_ref), 1e-30)
        assert np.all(np.abs(y_gpu - y_ref) <= 1e-5 * denom), "fp32 outputs differ by more than 1e-5 relative"
        assert np.array_equal(y_gpu, y_ref), "fp32 outputs are within tolerance but not identical"


def run_gemm_both(nq, case, x, full, **epi_kw):
    M = x.shape[0]
    out_int8 = epi_kw.get("out_int8", False)
    acc_ref = oracle.gemm_acc(x, case.ow_full if full else case.ow_part)
    y_ref = None
    dx = dev(x)
    fn = nq.nq_gemm_full if full else nq.nq_gemm_part
    for dump in (True, False):
        for kernel in each_kernel():
            epi, keep, okw = epi_pair(nq, case, full, (M,), dump=dump, **epi_kw)
            if y_ref is None:
                y_ref = oracle.epilogue(acc_ref, **okw)
            y = torch.full((M, case.N), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
            fn(dx, M, case.W.desc, epi, y)
            torch.cuda.synchronize()
            try:
                check_outputs(host(y), host(keep["acc"]) if dump else None, y_ref, acc_ref, out_int8)
            except AssertionError as e:
                raise AssertionError(f"{e} (kernel choice '{kernel}', accumulator dump {dump})") from None


def run_conv_both(nq, case, x, shape, full, **epi_kw):
    B, H, W, Cin = x.shape
    KH, KW, stride, pad = shape
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, stride, pad)
    out_int8 = epi_kw.get("out_int8", False)
    cs = nq.nq_conv_shape(B, H, W, Cin, case.N, KH, KW, stride, pad)
    fn = nq.nq_conv_full if full else nq.nq_conv_part
    w4 = (case.ow_full if full else case.ow_part).reshape(case.N, KH, KW, Cin)
    acc_ref = oracle.conv_acc(x, w4, stride, pad)
    y_ref = None
    dx = dev(x)
    for dump in (True, False):
        for kernel in each_kernel():
            epi, keep, okw = epi_pair(nq, case, full, (B, Ho, Wo), dump=dump, **epi_kw)
            if y_ref is None:
                y_ref = oracle.epilogue(acc_ref, **okw)
            y = torch.full((B, Ho, Wo, case.N), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
            fn(dx, cs, case.W.desc, epi, y)
            torch.cuda.synchronize()
            try:
                check_outputs(host(y), host(keep["acc"]) if dump else None, y_ref, acc_ref, out_int8)
            except AssertionError as e:
                raise AssertionError(f"{e} (kernel choice '{kernel}', accumulator dump {dump})") from None


def run_gconv_both(nq, case, x, shape, groups, full, **epi_kw):
    """Depthwise / grouped convolution: case holds [Cout, KH*KW*gs] weights, k = (kh*KW + kw)*gs + ci, gs = Cin / groups
    (Cout = case.N need not equal Cin)."""
    B, H, W, Cin = x.shape
    KH, KW, stride, pad = shape
    gs = Cin // groups
    C = case.N
    Ho, Wo = oracle.conv_out_hw(H, W, KH, KW, stride, pad)
    out_int8 = epi_kw.get("out_int8", False)
    cs = nq.nq_conv_shape(B, H, W, Cin, C, KH, KW, stride, pad)
    fn = nq.nq_gconv_full if full else nq.nq_gconv_part
    w4 = (case.ow_full if full else case.ow_part).reshape(C, KH, KW, gs)
    acc_ref = oracle.conv_grouped_acc(x, w4, groups, stride, pad)
    y_ref = None
    dx = dev(x)
    for dump in (True, False):
        epi, keep, okw = epi_pair(nq, case, full, (B, Ho, Wo), dump=dump, **epi_kw)
        if y_ref is None:
            y_ref = oracle.epilogue(acc_ref, **okw)
        y = torch.full((B, Ho, Wo, C), 77, dtype=torch.int8 if out_int8 else torch.float32, device="cuda")
        fn(dx, cs, groups, case.W.desc, epi, y)
        torch.cuda.synchronize()
        try:
            check_outputs(host(y), host(keep["acc"]) if dump else None, y_ref, acc_ref, out_int8)
        except AssertionError as e:
            raise AssertionError(f"{e} (accumulator dump {dump})") from None


from oracle.nq_oracle_cnn import oracle_cnn_forward  # noqa: E402,F401  (re-exported for the network tests)
