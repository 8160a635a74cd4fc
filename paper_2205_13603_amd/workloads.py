"""The workload table: for every named workload the operator, the instances of one device-filling launch, the
seeded synthetic inputs, the output shape and the roofline that bounds it.  Shared by the benchmark, the tuning
command and the tests.  No operator arithmetic and nothing of the CPU oracle lives here."""
from . import binding as B

# name -> (op factory, instances of one device-filling launch)
WORKLOADS = {
    "c1_gemm_f32_128": (lambda: B.gemm_op(128, 128, 128, "f32"), 4096),
    "c2_gemm_f16_1024": (lambda: B.gemm_op(1024, 1024, 1024, "f16"), 64),
    "x2_gemm_f8_1024": (lambda: B.gemm_op(1024, 1024, 1024, "f8", "f16"), 64),
    "c3_conv_f16_56x56x64": (lambda: B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1), 512),
    "c4a_bmm_nt_f16": (lambda: B.bmm_op(12, 128, 128, 64, True, "f16"), 1024),
    "c4b_bmm_nn_f16": (lambda: B.bmm_op(12, 128, 64, 128, False, "f16"), 1024),
    "c4c_gemm_i8_512": (lambda: B.gemm_op(512, 512, 512, "i8"), 512),
    "c5a_dw_f32_112x112x32": (lambda: B.dwconv2d_op(1, 112, 112, 32, stride=1, pad=1), 512),
    "c5b_dw_f32_56x56x144": (lambda: B.dwconv2d_op(1, 56, 56, 144, stride=2, pad=1), 512),
    "x5_cbr_f16_224x224x3": (lambda: B.conv2d_op(1, 224, 224, 3, 64, 7, 7, stride=2, pad=3), 256),
    "x5b_cbr_f16_224x224x4": (lambda: B.conv2d_op(1, 224, 224, 4, 64, 7, 7, stride=2, pad=3), 256),
    "x6_t2d_f16_4x4x512": (lambda: B.conv2d_transposed_op(1, 4, 4, 512, 256, 4, 4, stride=2, pad=1), 128),
    "x7_grp_f16_56x56x64_g4": (lambda: B.conv2d_op(1, 56, 56, 64, 128, 3, 3, stride=2, pad=1, groups=4), 512),
    "x8_gemm_nt_f16_1024": (lambda: B.bmm_op(1, 1024, 1024, 1024, True, "f16"), 64),
    "x9_c1d_f16_256x64": (lambda: B.conv1d_op(1, 256, 64, 128, 3, stride=2, pad=1), 4096),
    "x10_c3d_f16_16x224x224x3": (lambda: B.conv3d_op(1, 16, 224, 224, 3, 64, 7, stride=2, pad=3), 8),
    "x10b_c3d_f16_16x224x224x4": (lambda: B.conv3d_op(1, 16, 224, 224, 4, 64, 7, stride=2, pad=3), 8),
    "x11_gemm_bf16_1024": (lambda: B.gemm_op(1024, 1024, 1024, "bf16"), 64),
    "x12_conv_bf16_56x56x64": (lambda: B.conv2d_op(1, 56, 56, 64, 64, 3, 3, stride=1, pad=1, in_dtype="bf16"), 512),
    "x3_softmax_f32_256x256": (lambda: B.softmax_op(1, 256, 256), 2048),
    "x4_norm_f32_256x256": (lambda: B.norm_op(1, 256, 256), 2048),
}



def workload_inputs(name, seed):
    from . import inputs as I
    return {
        "c1_gemm_f32_128": lambda: list(I.c1(seed)),
        "c2_gemm_f16_1024": lambda: list(I.c2(seed)),
        "x2_gemm_f8_1024": lambda: list(I.c2(seed, dtype="f8")),
        "c3_conv_f16_56x56x64": lambda: list(I.c3(seed)),
        "c4a_bmm_nt_f16": lambda: list(I.c4a(seed)),
        "c4b_bmm_nn_f16": lambda: list(I.c4b(seed)),
        "c4c_gemm_i8_512": lambda: list(I.c4c(seed)),
        "c5a_dw_f32_112x112x32": lambda: list(I.c5a(seed)),
        "c5b_dw_f32_56x56x144": lambda: list(I.c5b(seed)),
        "x8_gemm_nt_f16_1024": lambda: list(I.c2nt(seed)),
        "x6_t2d_f16_4x4x512": lambda: list(I.t2d(seed)),
        "x9_c1d_f16_256x64": lambda: list(I.c1d(seed)),
        "x10_c3d_f16_16x224x224x3": lambda: list(I.c3d(seed)),
        "x10b_c3d_f16_16x224x224x4": lambda: list(I.c3d4(seed)),
        "x7_grp_f16_56x56x64_g4": lambda: list(I.grp(seed)),
        "x5_cbr_f16_224x224x3": lambda: list(I.cbr(seed)),
        "x5b_cbr_f16_224x224x4": lambda: list(I.cbr4(seed)),
        "x11_gemm_bf16_1024": lambda: list(I.c2(seed, dtype="bf16")),
        "x12_conv_bf16_56x56x64": lambda: list(I.c3(seed, dtype="bf16")),
        "x3_softmax_f32_256x256": lambda: list(I.sfm(seed)),
        "x4_norm_f32_256x256": lambda: list(I.nrm(seed)),
    }[name]()



OUT_SHAPE = {
    "c1_gemm_f32_128": ((128, 128), "f32"), "c2_gemm_f16_1024": ((1024, 1024), "f16"), "x2_gemm_f8_1024": ((1024, 1024), "f16"),
    "c3_conv_f16_56x56x64": ((1, 56, 56, 64), "f16"), "c4a_bmm_nt_f16": ((12, 128, 128), "f16"),
    "c4b_bmm_nn_f16": ((12, 128, 64), "f16"), "c4c_gemm_i8_512": ((512, 512), "i32"),
    "c5a_dw_f32_112x112x32": ((1, 112, 112, 32), "f32"), "c5b_dw_f32_56x56x144": ((1, 28, 28, 144), "f32"),
    "x3_softmax_f32_256x256": ((1, 256, 256), "f32"), "x4_norm_f32_256x256": ((1,), "f32"),
    "x5_cbr_f16_224x224x3": ((1, 112, 112, 64), "f16"), "x5b_cbr_f16_224x224x4": ((1, 112, 112, 64), "f16"),
    "x8_gemm_nt_f16_1024": ((1, 1024, 1024), "f16"), "x9_c1d_f16_256x64": ((1, 128, 128), "f16"),
    "x10_c3d_f16_16x224x224x3": ((1, 8, 112, 112, 64), "f16"), "x10b_c3d_f16_16x224x224x4": ((1, 8, 112, 112, 64), "f16"),
    "x11_gemm_bf16_1024": ((1024, 1024), "bf16"), "x12_conv_bf16_56x56x64": ((1, 56, 56, 64), "bf16"),
    "x6_t2d_f16_4x4x512": ((1, 8, 8, 256), "f16"), "x7_grp_f16_56x56x64_g4": ((1, 28, 28, 128), "f16"),
}
BOUND = {  # which roofline bounds the workload (AI vs ridge), and the in-dtype
    "c1_gemm_f32_128": ("alu", "f32"), "c2_gemm_f16_1024": ("mfma", "f16"), "c3_conv_f16_56x56x64": ("mfma", "f16"),
    "c4a_bmm_nt_f16": ("hbm", "f16"), "c4b_bmm_nn_f16": ("hbm", "f16"), "c4c_gemm_i8_512": ("hbm", "i8"),
    "c5a_dw_f32_112x112x32": ("hbm", "f32"), "c5b_dw_f32_56x56x144": ("hbm", "f32"),
    "x2_gemm_f8_1024": ("mfma", "f8"),  # beyond the eight configs: config 2 with 8-bit float inputs
    "x3_softmax_f32_256x256": ("hbm", "f32"), "x4_norm_f32_256x256": ("hbm", "f32"),  # row reductions
    "x5_cbr_f16_224x224x3": ("hbm", "f16"), "x5b_cbr_f16_224x224x4": ("hbm", "f16"),  # 122 flop per byte: below the ridge of 312
    "x7_grp_f16_56x56x64_g4": ("hbm", "f16"),  # 45 flop per byte
    "x8_gemm_nt_f16_1024": ("mfma", "f16"),  # config 2 with B stored [N][K] (both operands contiguous along k)
    "x9_c1d_f16_256x64": ("hbm", "f16"),  # 55 flop per byte
    "x10_c3d_f16_16x224x224x3": ("mfma", "f16"),  # 743 flop per byte
    "x10b_c3d_f16_16x224x224x4": ("mfma", "f16"),
    "x11_gemm_bf16_1024": ("mfma", "bf16"), "x12_conv_bf16_56x56x64": ("mfma", "bf16"),  # configs 2 and 3 in bfloat16
    "x6_t2d_f16_4x4x512": ("hbm", "f16"),  # 16 flop per byte: the 4 MiB of weights are read once per instance
}


PROFILE_NAME = {"c1_gemm_f32_128": "gemm_alu_c1_gemm_f32_128", "c2_gemm_f16_1024": "gemm_mfma_c2_gemm_f16_1024",
                "c3_conv_f16_56x56x64": "gemm_mfma_c3_conv_f16_56x56x64", "c5a_dw_f32_112x112x32": "dwconv_c5a_dw_f32_112x112x32",
                "c5b_dw_f32_56x56x144": "dwconv_c5b_dw_f32_56x56x144", "c4a_bmm_nt_f16": "gemm_mfma_c4a_bmm_nt_f16", "c4b_bmm_nn_f16": "gemm_mfma_c4b_bmm_nn_f16",
                "c4c_gemm_i8_512": "gemm_mfma_c4c_gemm_i8_512", "x2_gemm_f8_1024": "gemm_mfma_x2_gemm_f8_1024",
                "x3_softmax_f32_256x256": "reduce_x3_softmax_f32_256x256", "x4_norm_f32_256x256": "reduce_x4_norm_f32_256x256",
                "x5_cbr_f16_224x224x3": "gemm_mfma_x5_cbr_f16_224x224x3", "x5b_cbr_f16_224x224x4": "gemm_mfma_x5b_cbr_f16_224x224x4",
                "x10_c3d_f16_16x224x224x3": "gemm_mfma_x10_c3d_f16_16x224x224x3", "x10b_c3d_f16_16x224x224x4": "gemm_mfma_x10b_c3d_f16_16x224x224x4", "x6_t2d_f16_4x4x512": "gemm_mfma_x6_t2d_f16_4x4x512",
                "x7_grp_f16_56x56x64_g4": "gemm_mfma_x7_grp_f16_56x56x64_g4", "x8_gemm_nt_f16_1024": "gemm_mfma_x8_gemm_nt_f16_1024",
                "x9_c1d_f16_256x64": "gemm_mfma_x9_c1d_f16_256x64", "x11_gemm_bf16_1024": "gemm_mfma_x11_gemm_bf16_1024",
                "x12_conv_bf16_56x56x64": "gemm_mfma_x12_conv_bf16_56x56x64"}
