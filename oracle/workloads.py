"""The oracle's result for one instance of a named workload (test infrastructure: used by the GPU parity
tests, by bench.py's correctness check and by its cpu_baseline leg; the product never imports this)."""
from . import oracle as O


def oracle_run(name, ins):
    if name in ("c1_gemm_f32_128", "c2_gemm_f16_1024", "c4c_gemm_i8_512", "x2_gemm_f8_1024"):
        return O.gemm(ins[0], ins[1])
    if name == "x11_gemm_bf16_1024":
        return O.gemm(ins[0], ins[1], bf16=True)
    if name == "x12_conv_bf16_56x56x64":
        return O.conv2d_nhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=1, pad=1, bf16=True)
    if name == "c4a_bmm_nt_f16":
        return O.bmm(ins[0], ins[1], trans_b=True)
    if name == "c4b_bmm_nn_f16":
        return O.bmm(ins[0], ins[1])
    if name == "c3_conv_f16_56x56x64":
        return O.conv2d_nhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=1, pad=1)
    if name == "c5a_dw_f32_112x112x32":
        return O.dwconv2d_nhwc(ins[0], ins[1], stride=1, pad=1)
    if name == "c5b_dw_f32_56x56x144":
        return O.dwconv2d_nhwc(ins[0], ins[1], stride=2, pad=1)
    if name == "x7_grp_f16_56x56x64_g4":
        return O.conv2d_nhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=2, pad=1, groups=4)
    if name == "x8_gemm_nt_f16_1024":
        return O.bmm(ins[0], ins[1], trans_b=True)
    if name in ("x10_c3d_f16_16x224x224x3", "x10b_c3d_f16_16x224x224x4"):
        return O.conv3d_ndhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=2, pad=3)
    if name == "x9_c1d_f16_256x64":
        return O.conv1d_nwc(ins[0], ins[1], bias=ins[2], relu=True, stride=2, pad=1)
    if name == "x6_t2d_f16_4x4x512":
        return O.conv2d_transposed_nhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=2, pad=1)
    if name in ("x5_cbr_f16_224x224x3", "x5b_cbr_f16_224x224x4"):
        return O.conv2d_nhwc(ins[0], ins[1], bias=ins[2], relu=True, stride=2, pad=3)
    if name == "x3_softmax_f32_256x256":
        return O.softmax(ins[0])
    if name == "x4_norm_f32_256x256":
        return O.norm(ins[0])
    raise KeyError(name)
