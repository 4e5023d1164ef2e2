"""Small layers for GPU parity: every shape spans several kernel tiles and ends in a ragged tail."""
import vq_synth as s

# name -> make_layer keyword arguments (config id 300+ keeps their seeds apart from the benchmark layers)
SMALL = {
    "v6_k256": dict(out_features=70, in_features=391, v=6, k=256),
    "v6_k4096": dict(out_features=261, in_features=1030, v=6, k=4096),
    "v6_k4096_res4096": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096),
    "v6_res256_outlier": dict(out_features=150, in_features=1207, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096),
    "v8_k65536": dict(out_features=200, in_features=520, v=8, k=65536),
    "v8_fused_path": dict(out_features=200, in_features=768, v=8, k=65536),                # in % 256 == 0: the fused MFMA kernel
    "v8_k256": dict(out_features=131, in_features=2056, v=8, k=256),                         # 8-bit indices; 257 vectors: one past a step of 256
    "v8_k65536_res256": dict(out_features=203, in_features=4096, v=8, k=65536, k_res=256),   # the residual setting of the 2-bit tables
    "v8_long_rows": dict(out_features=203, in_features=8200, v=8, k=65536, k_res=256),        # from 8192 columns on a wave takes two rows (203: a last wave with one)
    "v8_k65536_res65536": dict(out_features=77, in_features=1536, v=8, k=65536, k_res=65536),
    "v8_k200_res40000": dict(out_features=2050, in_features=264, v=8, k=200, k_res=40000, with_scale=False),
    "v8_k65536_unscaled": dict(out_features=129, in_features=264, v=8, k=65536, with_scale=False, with_bias=False),
    "odd_everything": dict(out_features=37, in_features=203, v=5, k=37, k_res=11, n_outlier_cols=9, v_out=3, k_out=5),
    "v1_k2": dict(out_features=9, in_features=77, v=1, k=2),
    "v16_k300": dict(out_features=33, in_features=530, v=16, k=300, with_scale=False),
    "v2_k16_nobias": dict(out_features=65, in_features=130, v=2, k=16, with_bias=False),
    "v4_k256_res16": dict(out_features=64, in_features=256, v=4, k=256, k_res=16),
    "v12_k4096_res4096": dict(out_features=40, in_features=600, v=12, k=4096, k_res=4096),
    "single_row": dict(out_features=1, in_features=4096, v=6, k=4096),
    "single_vector": dict(out_features=300, in_features=5, v=6, k=4096),
    "v6_exact_fit": dict(out_features=3, in_features=6144, v=6, k=4096, k_res=4096),      # stream fills its row stride exactly
    "v6_many_rows": dict(out_features=9000, in_features=390, v=6, k=4096, k_res=256),    # several row chunks per workgroup
    "v6_wide_outlier": dict(out_features=70, in_features=2600, v=6, k=4096, n_outlier_cols=1200, v_out=4, k_out=4096),
    "padded_stride": dict(out_features=50, in_features=300, v=6, k=4096, k_res=256, extra_stride=2),
    # the matrix-core GEMV: more 16-row blocks per workgroup than one chunk holds (4, 3 or 2 by residual kind), a ragged
    # last block, and more column passes per wave than its prefetch ring holds
    "v6_chunks": dict(out_features=20501, in_features=198, v=6, k=4096),
    "v6_chunks_res8_outlier": dict(out_features=16421, in_features=210, v=6, k=4096, k_res=256, n_outlier_cols=12, v_out=4, k_out=4096),
    "v6_chunks_res12": dict(out_features=12303, in_features=198, v=6, k=4096, k_res=4096),
    "v6_passes": dict(out_features=40, in_features=7000, v=6, k=4096, k_res=4096),
    "v6_passes_res8": dict(out_features=37, in_features=9100, v=6, k=4096, k_res=256),
    # tables shorter than their index widths allow (the one-row kernel for 8-bit residual streams clamps its table loads), an
    # outlier table in the padding of the other two, more rows than one round of its ring
    "v6_short_tables_res8_outlier": dict(out_features=2300, in_features=2500, v=6, k=3000, k_res=200, n_outlier_cols=40, v_out=4, k_out=2100),
    # in_features a multiple of 256: vq_gemm's restore-then-multiply route (with a workspace) takes any layer
    "v6_dense_gemm": dict(out_features=203, in_features=1024, v=6, k=4096, k_res=4096, n_outlier_cols=16, v_out=4, k_out=4096),
    # codebook groups: a table (and residual table) per range of vectors.  Group sizes that are multiples of 8 vectors run
    # on the fast kernels (ragged last group, groups narrower than one pass of the eight waves, several chunks of rows
    # whose sums wait in LDS for the next group, groups longer than the prefetch ring); the others on the generic ones
    "grp_v6": dict(out_features=261, in_features=1030, v=6, k=4096, group_vectors=64),
    "grp_v6_res12": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096, group_vectors=40),
    "grp_v6_res8_outlier": dict(out_features=150, in_features=1207, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096, group_vectors=64),
    "grp_v6_chunks": dict(out_features=20501, in_features=198, v=6, k=4096, group_vectors=16),
    "grp_v6_chunks_res12": dict(out_features=12303, in_features=390, v=6, k=4096, k_res=4096, group_vectors=24),
    "grp_v6_passes": dict(out_features=40, in_features=7000, v=6, k=4096, k_res=4096, group_vectors=600),
    "grp_v6_sixteen": dict(out_features=300, in_features=4096, v=6, k=4096, group_vectors=48),
    "grp_v6_narrow_res8": dict(out_features=3000, in_features=1150, v=6, k=4096, k_res=256, group_vectors=32),
    "grp_v6_small_tables": dict(out_features=70, in_features=391, v=6, k=3000, k_res=200, group_vectors=8),
    "grp_v6_unaligned": dict(out_features=70, in_features=800, v=6, k=4096, k_res=256, group_vectors=20),
    "v6_res12_outliers_tall": dict(out_features=2500, in_features=1136, v=6, k=4096, k_res=4096, n_outlier_cols=136, v_out=4, k_out=300),   # outlier table left in global memory
    "grp_v6_dense_gemm": dict(out_features=203, in_features=1024, v=6, k=4096, k_res=4096, n_outlier_cols=16, v_out=4, k_out=4096, group_vectors=56),
    "grp_v8": dict(out_features=200, in_features=768, v=8, k=65536, group_vectors=40),
    "grp_odd": dict(out_features=37, in_features=203, v=5, k=37, k_res=11, n_outlier_cols=9, v_out=3, k_out=5, group_vectors=7),
    # vectors down the output dimension (the paper's orientation): rows not a multiple of v, outlier columns not a multiple
    # of v_out, codebook groups over columns, a big table
    "down_v6": dict(out_features=70, in_features=391, v=6, k=4096, orientation=1),
    "down_v6_res_outlier": dict(out_features=150, in_features=1207, v=6, k=4096, k_res=256, n_outlier_cols=25, v_out=4, k_out=4096, orientation=1),
    "down_v8_k65536": dict(out_features=200, in_features=520, v=8, k=65536, orientation=1),
    "down_v8_k256_res65536": dict(out_features=203, in_features=1100, v=8, k=256, k_res=65536, orientation=1),   # a ragged last stream; one wave without columns
    "down_v8_outliers": dict(out_features=100, in_features=612, v=8, k=65536, k_res=256, n_outlier_cols=12, v_out=4, k_out=16, orientation=1),
    "down_v8_groups_res256": dict(out_features=64, in_features=3001, v=8, k=65536, k_res=256, group_vectors=300, orientation=1, with_bias=False),
    "down_groups": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096, group_vectors=100, orientation=1),
    "down_odd": dict(out_features=37, in_features=203, v=5, k=37, k_res=11, n_outlier_cols=9, v_out=3, k_out=5, orientation=1),
    "down_v16": dict(out_features=33, in_features=530, v=16, k=300, with_scale=False, orientation=1),
    # ... and the shapes of the fast kernel for that orientation (v = 6, 12-bit indices, no outlier columns, rows of x on
    # 16-byte boundaries): ragged last stream and last pass, more stream groups than workgroups, streams split over waves
    "down_fast_v6": dict(out_features=70, in_features=392, v=6, k=4096, orientation=1),
    "down_fast_res12": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096, orientation=1),
    "down_fast_res8": dict(out_features=150, in_features=1208, v=6, k=4096, k_res=256, orientation=1),
    "down_fast_many_streams": dict(out_features=20501, in_features=200, v=6, k=4096, orientation=1),
    "down_fast_long": dict(out_features=40, in_features=7000, v=6, k=4096, k_res=4096, orientation=1),
    "down_fast_small_tables": dict(out_features=300, in_features=4096, v=6, k=3000, k_res=200, with_bias=False, orientation=1),
    "down_fast_outlier": dict(out_features=150, in_features=1208, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096, orientation=1),
    "down_fast_outlier_41": dict(out_features=261, in_features=2040, v=6, k=4096, n_outlier_cols=41, v_out=4, k_out=4096, orientation=1),
    "down_fast_outlier_many_streams": dict(out_features=20501, in_features=208, v=6, k=4096, k_res=4096, n_outlier_cols=70, v_out=5, k_out=300, orientation=1),
    "down_fast_parts": dict(out_features=1000, in_features=2104, v=6, k=4096, k_res=4096, orientation=1),
    # ... with codebook groups over the columns (fast only with a workspace: tests of vq_gemv_with_workspace)
    "down_fast_groups": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096, group_vectors=104, orientation=1),
    "down_fast_groups_outlier": dict(out_features=150, in_features=1208, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096,
                                     group_vectors=200, orientation=1),
    "down_fast_groups_outlier_tall": dict(out_features=5003, in_features=1240, v=6, k=4096, k_res=4096, n_outlier_cols=40, v_out=8,
                                          k_out=300, group_vectors=200, orientation=1),
    "down_fast_long_rows_res12": dict(out_features=66, in_features=16000, v=6, k=4096, k_res=4096, orientation=1),
    "down_fast_groups_many": dict(out_features=5000, in_features=4096, v=6, k=4096, group_vectors=600, orientation=1),
    "down_dense_gemm": dict(out_features=203, in_features=1024, v=6, k=4096, k_res=4096, n_outlier_cols=16, v_out=4, k_out=4096, orientation=1),
    # the paper's other (v, k) settings on the decode kernels that keep the tables in LDS: whole-window index loads for
    # 4-, 8- and 12-bit streams (ragged last window, rows past a multiple of sixteen, a residual stream of the same width, a
    # permutation), and the run-time variant for everything else (residual of another width, outlier columns)
    "lds_v4_k256": dict(out_features=517, in_features=1030, v=4, k=256),
    "lds_v4_k256_res256": dict(out_features=300, in_features=2052, v=4, k=256, k_res=256),
    "lds_v2_k16": dict(out_features=1000, in_features=650, v=2, k=16, with_scale=False),
    "lds_v12_k4096": dict(out_features=77, in_features=3000, v=12, k=4096),
    "lds_v8_k4096": dict(out_features=260, in_features=1000, v=8, k=3000, k_res=4000),
    "lds_v4_k4096_perm": dict(out_features=130, in_features=1023, v=4, k=4096, permute=True),
    "lds_v4_k256_outlier": dict(out_features=130, in_features=1030, v=4, k=256, k_res=16, n_outlier_cols=16, v_out=2, k_out=64),
    # two tables that do not fit LDS together (v = 12 with two 4096-entry tables: Table "Quantization parameters", the 2.26-bit
    # setting): one table at a time, two passes over the rows; several rows per wave; long rows of v = 8
    "lds_v12_two_tables": dict(out_features=5000, in_features=1500, v=12, k=4096, k_res=4096),
    "lds_v12_two_tables_perm": dict(out_features=77, in_features=3001, v=12, k=4000, k_res=3000, permute=True, with_bias=False),
    "lds_v8_two_tables_long": dict(out_features=100, in_features=20000, v=8, k=4096, k_res=4096),
    # the 2.07- to 2.26-bit settings of that table: codebook groups (not in whole windows), 1 % outlier columns of v = 4 with
    # 8192 entries (13 index bits), a permutation; one table in LDS per pass
    "lds_v12_groups_res_outlier": dict(out_features=300, in_features=2000, v=12, k=4096, k_res=4096, n_outlier_cols=20, v_out=4,
                                       k_out=8192, group_vectors=50),
    "lds_v12_groups_perm": dict(out_features=5000, in_features=1500, v=12, k=4000, k_res=3000, group_vectors=40, permute=True),
    "lds_v4_k256_groups": dict(out_features=517, in_features=1030, v=4, k=256, k_res=256, group_vectors=100),
    "lds_v6_outlier13": dict(out_features=150, in_features=1208, v=6, k=4096, n_outlier_cols=24, v_out=4, k_out=8192),
    "lds_v12_outlier_only": dict(out_features=130, in_features=1500, v=12, k=4096, n_outlier_cols=16, v_out=4, k_out=4096, with_scale=False),
    # ... and the same settings stored with vectors down the output dimension (Sec. 3.1): streams of v rows, a ragged last
    # stream, outlier streams of 4 rows (also under v = 6 streams), groups of columns, a permutation
    "down_lds_v12_two_tables": dict(out_features=1000, in_features=900, v=12, k=4096, k_res=4096, orientation=1),
    "down_lds_v12_groups_outlier": dict(out_features=530, in_features=1200, v=12, k=4000, k_res=3000, n_outlier_cols=12, v_out=4, k_out=8192,
                                        group_vectors=300, orientation=1),
    "down_lds_v4_k256_perm": dict(out_features=203, in_features=2000, v=4, k=256, k_res=256, orientation=1, permute=True),
    "down_lds_v6_outlier13": dict(out_features=151, in_features=700, v=6, k=4096, n_outlier_cols=21, v_out=4, k_out=8192, orientation=1),
    "down_lds_v2_k16": dict(out_features=77, in_features=3000, v=2, k=16, orientation=1, with_bias=False),
    "down_lds_v12_odd_groups": dict(out_features=100, in_features=1001, v=12, k=4096, k_res=4096, group_vectors=333, orientation=1),
    "down_lds_v8_many_streams": dict(out_features=30011, in_features=300, v=8, k=4096, k_res=3000, orientation=1),
    # vq_gemm's on-the-fly kernel for v = 6 (tables in LDS; in_features a multiple of 256, no outlier columns, one group):
    # no residual, 8-bit and 12-bit residual streams, short tables, a ragged last channel block
    "v6_gemm_plain": dict(out_features=300, in_features=768, v=6, k=4096),
    "v6_gemm_res8": dict(out_features=200, in_features=512, v=6, k=3000, k_res=200),
    "v6_gemm_res12": dict(out_features=133, in_features=1024, v=6, k=4096, k_res=4096, with_bias=False),
    # ... with outlier columns in whole runs of 16 (a whole step, a step and a half, half a step; a ragged last main vector)
    "v6_gemm_outlier32": dict(out_features=200, in_features=512, v=6, k=4096, k_res=256, n_outlier_cols=32, v_out=4, k_out=4096),
    "v6_gemm_outlier48": dict(out_features=133, in_features=768, v=6, k=3000, n_outlier_cols=48, v_out=3, k_out=100),
    "v6_gemm_outlier16_res12": dict(out_features=140, in_features=512, v=6, k=4096, k_res=4096, n_outlier_cols=16, v_out=2, k_out=16),
    # stored column order a permutation of the layer's (the outlier columns scattered over the layer): the kernels that
    # gather the activations themselves, the generic ones, both orientations, groups, the long-row kernel, both vq_gemm routes
    "perm_v6_k4096": dict(out_features=261, in_features=1030, v=6, k=4096, permute=True),
    "perm_v6_res12": dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096, permute=True),
    "perm_v6_res8_outlier": dict(out_features=150, in_features=1208, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096, permute=True),
    "perm_v6_res8_outlier_odd": dict(out_features=150, in_features=1207, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096, permute=True),
    "perm_v6_long_res8_outlier": dict(out_features=300, in_features=16400, v=6, k=4096, k_res=256, n_outlier_cols=40, v_out=4, k_out=4096, permute=True),
    "perm_v6_dense_gemm": dict(out_features=203, in_features=1024, v=6, k=4096, k_res=4096, n_outlier_cols=16, v_out=4, k_out=4096, permute=True),
    "perm_grp_v6": dict(out_features=261, in_features=1030, v=6, k=4096, group_vectors=64, permute=True),
    "perm_v8_fused_path": dict(out_features=200, in_features=768, v=8, k=65536, permute=True),
    "perm_odd": dict(out_features=37, in_features=203, v=5, k=37, k_res=11, n_outlier_cols=9, v_out=3, k_out=5, permute=True),
    "perm_down_fast_outlier": dict(out_features=150, in_features=1208, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096, orientation=1, permute=True),
    "perm_down_v8": dict(out_features=200, in_features=520, v=8, k=65536, orientation=1, permute=True),
}


def small_layer(name):
    kw = dict(SMALL[name])
    return s.make_layer(300 + list(SMALL).index(name), name, kw.pop("out_features"), kw.pop("in_features"),
                        kw.pop("v"), kw.pop("k"), **kw)


# Sets of layers that read the same activations, for vq_gemv_multi: name -> list of make_layer keyword arguments.
MULTI = {
    "qkv_v6": [dict(out_features=261, in_features=1030, v=6, k=4096), dict(out_features=70, in_features=1030, v=6, k=4096),
               dict(out_features=133, in_features=1030, v=6, k=3000)],
    "gate_up_res12": [dict(out_features=133, in_features=1000, v=6, k=4096, k_res=4096),
                      dict(out_features=150, in_features=1000, v=6, k=4096, k_res=4096, with_bias=False)],
    "res8_outlier_pair": [dict(out_features=150, in_features=1207, v=6, k=4096, k_res=256, n_outlier_cols=24, v_out=4, k_out=4096),
                          dict(out_features=47, in_features=1207, v=6, k=4096, k_res=256)],
    # many 16-row blocks per workgroup, different for each layer, ragged last blocks
    "many_rows": [dict(out_features=20501, in_features=198, v=6, k=4096), dict(out_features=12303, in_features=198, v=6, k=4096),
                  dict(out_features=5, in_features=198, v=6, k=4096)],
    "eight_layers": [dict(out_features=40 + 16 * i, in_features=600, v=6, k=4096, k_res=256) for i in range(8)],
    # sets that the fused kernel does not take together: they run one after the other
    "mixed_residual_kinds": [dict(out_features=70, in_features=1000, v=6, k=4096), dict(out_features=70, in_features=1000, v=6, k=4096, k_res=4096)],
    "with_groups": [dict(out_features=70, in_features=1000, v=6, k=4096, group_vectors=64), dict(out_features=33, in_features=1000, v=6, k=4096)],
    "generic_shapes": [dict(out_features=200, in_features=520, v=8, k=65536), dict(out_features=37, in_features=520, v=5, k=37, k_res=11)],
    "single": [dict(out_features=261, in_features=1030, v=6, k=4096)],
    # layers with vectors down the output dimension: one launch of that orientation's matrix-core kernel for any batch
    "down_qkv": [dict(out_features=261, in_features=1032, v=6, k=4096, orientation=1), dict(out_features=70, in_features=1032, v=6, k=4096, orientation=1),
                 dict(out_features=133, in_features=1032, v=6, k=3000, orientation=1)],
    "down_gate_up_res12_outlier": [dict(out_features=133, in_features=1208, v=6, k=4096, k_res=4096, orientation=1),
                                   dict(out_features=1150, in_features=1208, v=6, k=4096, k_res=4096, n_outlier_cols=24, v_out=4, k_out=4096,
                                        with_bias=False, orientation=1)],
    "down_res8_many_streams": [dict(out_features=20501, in_features=200, v=6, k=4096, k_res=256, orientation=1),
                               dict(out_features=5, in_features=200, v=6, k=4096, k_res=256, orientation=1)],
    # ... and sets that run one after the other: both orientations, codebook groups
    "down_and_rowwise": [dict(out_features=70, in_features=1000, v=6, k=4096, orientation=1), dict(out_features=70, in_features=1000, v=6, k=4096)],
    "down_with_groups": [dict(out_features=70, in_features=1000, v=6, k=4096, group_vectors=64, orientation=1),
                         dict(out_features=33, in_features=1000, v=6, k=4096, orientation=1)],
}


def multi_layers(name):
    out = []
    for i, kw in enumerate(MULTI[name]):
        kw = dict(kw)
        out.append(s.make_layer(400 + list(MULTI).index(name), "%s_%d" % (name, i), kw.pop("out_features"), kw.pop("in_features"),
                                kw.pop("v"), kw.pop("k"), layer_ordinal=i, **kw))
    return out
