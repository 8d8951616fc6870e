"""The labels the profile summaries give to this library's kernels (rocprofv3 prints long names mangled and short
ones demangled): the two kernels of a forward pass, the sweep and the layout pre-passes must stay distinguishable."""
from paper_2507_07966_amd.profile_summary import short_name

PASS = "_ZN2pa12_GLOBAL__N_116pass_bf16_kernelILi128ELb%dELi%dELb%dELb%dEEEvPKDF16bS3_S3_PfS4_PKfS6_PDF16bS4_PKNS_8WorkItemE"


def test_forward_pass_labels():
    assert short_name(PASS % (0, 0, 0, 0)) == "prefix_pass (bf16 MFMA)"
    assert short_name(PASS % (0, 0, 0, 1)) == "careful kernel of the prefix pass"
    assert short_name(PASS % (1, 1, 1, 0)) == "attention_sweep (bf16 MFMA)"
    assert short_name(PASS % (1, 0, 1, 0)) == "attention_sweep (bf16 MFMA), fp32 partial"
    assert short_name(PASS % (1, 1, 1, 1)) == "careful kernel of the sweep"
    assert short_name(PASS % (1, 2, 0, 0)) == "suffix_pass (bf16 MFMA), merging"
    assert short_name(PASS % (1, 1, 0, 0)) == "suffix_pass (bf16 MFMA), final"
    assert short_name(PASS % (1, 0, 0, 1)) == "careful kernel of the suffix pass"
    # a label that starts with the common kernel's name would be summed into it by the profile scripts
    for causal, epi, sweep in ((0, 0, 0), (1, 1, 1), (1, 2, 0)):
        common, careful = short_name(PASS % (causal, epi, sweep, 0)), short_name(PASS % (causal, epi, sweep, 1))
        assert not careful.startswith(common.split(" (")[0])


def test_layout_prepass_labels():
    v = "void pa::(anonymous namespace)::vt_image_kernel<128, false>(unsigned short const*, unsigned short const*)"
    k = "void pa::(anonymous namespace)::vt_image_kernel<128, true>(unsigned short const*, unsigned short const*)"
    assert short_name(v) == "v_layout_prepass" and short_name(k) == "k_layout_prepass (backward)"
    assert short_name("_ZN2pa12_GLOBAL__N_115vt_image_kernelILi64ELb1EEEvPKtS3_PtS4_PKiS6_liiii") == "k_layout_prepass (backward)"
    assert short_name("_ZN2pa12_GLOBAL__N_115vt_image_kernelILi64ELb0EEEvPKtS3_PtS4_PKiS6_liiii") == "v_layout_prepass"


def test_other_kernel_labels():
    assert short_name("_ZN2pa12_GLOBAL__N_119logprob_tile_kernelEPKDF16bS2_PKiP15HIP_vector_typeIfLj2EEPfliiiiif").startswith("logprob_tile")
    assert short_name("_ZN2pa12_GLOBAL__N_114merge_n_kernelILi128EEEvPKPKfS5_") == "merge_partials (n-way)"
    assert short_name("_ZN2pa12_GLOBAL__N_113bwd_dq_kernelILi128ELb0EEEvPKDF16b") == "bwd_dq (bf16 MFMA)"
    assert short_name("_ZN2pa12_GLOBAL__N_113bwd_dq_kernelILi128ELb1EEEvPKDF16b") == "bwd_dq (bf16 MFMA), key splits"
