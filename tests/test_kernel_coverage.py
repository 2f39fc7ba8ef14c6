"""Every kernel instantiation compiled into libsparrow.so and the GPU test that runs it against the
oracle.  The table below is checked two ways on the CPU: its keys must be exactly the set of
`__global__` instantiations the library holds (read from the library's host stubs, so a new
template instance cannot appear without a line here), and every test it names must exist.  That
each line is true was observed with a kernel trace of every GPU test file
(profiles/gpu_test_suite_kernel_coverage.txt).

instantiation                                   test file : test (parameters)
"""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2602_15318_amd", "libsparrow.so")

A, AC, AS, ASQ, T, H, C, G = ("test_gpu_parity_attn.py", "test_gpu_parity_accept.py",
                              "test_gpu_parity_accept_sample.py", "test_gpu_parity_accept_sample_q.py",
                              "test_gpu_parity_tree.py", "test_gpu_parity_hsr.py",
                              "test_gpu_parity_commit.py", "test_gpu_graph_and_passes.py")

COVERAGE = {
    # ---- verification attention, matrix cores (bf16, d = 128): <steps in flight, row tiles>
    "verify_partial_mfma_kernel<1, 1>": (A, "test_c5_bf16_26k_chain8_layer", "C5 layer, C2; chains up to 64 rows per KV head"),
    "verify_partial_mfma_kernel<2, 1>": (A, "test_c4_bf16_ragged_batch8", "splits longer than 10 steps: ragged batch"),
    "verify_partial_mfma_kernel<1, 2>": (A, "test_paper_sized_trees_at_26k_context", "16-node tree: one block of 128 rows, short splits"),
    "verify_partial_mfma_kernel<2, 2>": (A, "test_c3_bf16_26k_tree60", "C3 60-node tree and the 30-node tree: blocks of 128 rows"),
    "verify_partial_mfma_kernel<1, 3>": (A, "test_paper_sized_trees_at_26k_context", "48-, 44- and 25-node trees: blocks of 192 rows"),
    "verify_combine_tiled_kernel<16>": (A, "test_c5_bf16_26k_chain8_layer", "more than 32 splits per sequence"),
    "verify_combine_tiled_kernel<8>": (A, "test_paper_sized_trees_at_26k_context", "17 to 32 splits (30-, 48-node trees)"),
    "verify_combine_tiled_kernel<4>": (A, "test_c3_bf16_26k_tree60", "at most 16 splits (C3, C4, batches)"),
    # ---- verification attention, plain ALU: <storage type, head_dim>
    "verify_partial_generic_kernel<float, 64>": (A, "test_c1_fp32", "C1"),
    "verify_combine_kernel<float, 64>": (A, "test_c1_fp32", "C1"),
    "verify_partial_generic_kernel<float, 128>": (A, "test_verify_context_lengths", "f32-8-2-128"),
    "verify_combine_kernel<float, 128>": (A, "test_verify_context_lengths", "f32-8-2-128"),
    "verify_partial_generic_kernel<unsigned short, 64>": (A, "test_verify_context_lengths", "bf16-8-2-64"),
    "verify_combine_kernel<unsigned short, 64>": (A, "test_verify_context_lengths", "bf16-8-2-64"),
    "verify_partial_generic_kernel<unsigned short, 128>": (A, "test_kv_span_of_2_gib_takes_the_plain_alu_kernels", "K/V span of 2 GiB"),
    "verify_combine_kernel<unsigned short, 128>": (A, "test_kv_span_of_2_gib_takes_the_plain_alu_kernels", "K/V span of 2 GiB"),
    # ---- draft window attention: <storage type, head_dim>
    "draft_window_attn_kernel<float, 64>": (A, "test_c1_fp32", "C1"),
    "draft_window_attn_kernel<float, 128>": (A, "test_draft_windows_and_layouts", "f32-8-2-128"),
    "draft_window_attn_kernel<unsigned short, 64>": (A, "test_draft_windows_and_layouts", "bf16-8-2-64"),
    "draft_window_attn_kernel<unsigned short, 128>": (A, "test_c2_bf16_8k_chain5", "C2 to C5"),
    # ---- lm_head + argmax + acceptance
    "lm_head_generic_kernel<float>": (AC, "test_c1_fp32_accept", "C1"),
    "lm_head_generic_kernel<unsigned short>": (AC, "test_accept_shapes", "bf16-520-777: hidden not a multiple of 512"),
    "lm_head_mfma_kernel": (AC, "test_accept_shapes", "bf16-512-4096, bf16-1024-9000"),
    "lm_head_ksplit_kernel<7, 1>": (AC, "test_c5_full_vocab_accept", "hidden 3584, at most 16 rows"),
    "lm_head_ksplit_kernel<7, 2>": (AC, "test_accept_shapes", "bf16-3584-8192-8-6 / 8-7: 17-32 rows and the paired 64-row pass"),
    "lm_head_ksplit_kernel<8, 1>": (AC, "test_accept_shapes", "bf16-4096-6000-1-8"),
    "lm_head_ksplit_kernel<8, 2>": (AC, "test_accept_shapes", "bf16-4096-6000-4-7, 3-10, 8-7"),
    "accept_finalize_kernel": (AC, "test_accept_shapes", "every greedy case"),
    "logit_stats_kernel": (AS, "test_accept_sample_matches_oracle", "every stochastic case"),
    "accept_sample_kernel": (AS, "test_accept_sample_matches_oracle", "deterministic children"),
    "accept_sample_q_kernel": (ASQ, "test_accept_sample_q_matches_oracle", "sampled draft"),
    # ---- dynamic draft tree
    "topk_chunk_kernel": (T, "test_draft_topk", ""),
    "topk_merge_kernel": (T, "test_draft_topk", ""),
    "tree_expand_kernel": (T, "test_tree_expand_and_select", ""),
    "tree_select_kernel": (T, "test_tree_expand_and_select", ""),
    # ---- draft input and post-accept commit
    "hsr_fc_generic_kernel<float>": (H, "test_hsr_fc", "f32-4-1-64-256"),
    "hsr_fc_generic_kernel<unsigned short>": (H, "test_hsr_fc", "bf16-4-2-64-512"),
    "hsr_fc_mfma_kernel<7, 2>": (H, "test_hsr_fc", "bf16-28-4-128-3584"),
    "hsr_fc_mfma_kernel<8, 2>": (H, "test_hsr_fc", "bf16-32-8-128-4096"),
    "hsr_fc_gemv_kernel<14>": (H, "test_hsr_fc", "bf16-28-4-128-3584, one row"),
    "hsr_fc_gemv_kernel<16>": (H, "test_hsr_fc", "bf16-32-8-128-4096, one row"),
    "draft_qkv_gemv_kernel<7>": (H, "test_draft_qkv_append", "bf16-28-4-128-3584, one row"),
    "draft_qkv_gemv_kernel<8>": (H, "test_draft_qkv_append", "bf16-32-8-128-4096, one row"),
    "draft_qkv_generic_kernel<float>": (H, "test_draft_qkv_append", "f32-4-1-64-256"),
    "draft_qkv_generic_kernel<unsigned short>": (H, "test_draft_qkv_append", "bf16-4-2-64-512"),
    "draft_qkv_mfma_kernel<7, 1>": (H, "test_draft_qkv_append", "bf16-28-4-128-3584"),
    "draft_qkv_mfma_kernel<8, 1>": (H, "test_draft_qkv_append", "bf16-32-8-128-4096"),
    "kv_commit_kernel": (C, "test_kv_commit_bit_exact", ""),
    # ---- measurement aid (no part of the method, nothing to compare): run, input left alone
    "stream_read_kernel<2>": (G, "test_stream_read_shapes_run", ""),
    "stream_read_kernel<4>": (G, "test_stream_read_shapes_run", ""),
    "stream_read_kernel<8>": (G, "test_stream_read_shapes_run", ""),
    "stream_read_kernel<16>": (G, "test_stream_read_shapes_run", ""),
}


def _compiled_instantiations():
    if not os.path.exists(LIB):
        from paper_2602_15318_amd import build
        build.build()
    out = subprocess.run(["nm", "-C", LIB], capture_output=True, text=True, check=True).stdout
    names = set()
    for line in out.splitlines():
        m = re.search(r"__device_stub__(.*?)\(", line)
        if m:
            names.add(m.group(1))
    return names


def test_every_compiled_kernel_instantiation_has_a_test():
    compiled = _compiled_instantiations()
    assert len(compiled) >= 40, "could not read the kernel list from the library"
    assert compiled == set(COVERAGE), (
        f"not in the table: {sorted(compiled - set(COVERAGE))}; in the table but not compiled: "
        f"{sorted(set(COVERAGE) - compiled)}")


def test_the_named_tests_exist():
    for kernel, (fname, test, _) in COVERAGE.items():
        src = open(os.path.join(ROOT, "tests", fname)).read()
        assert re.search(rf"^def {test}\(", src, flags=re.M), f"{kernel}: {fname} has no {test}"
