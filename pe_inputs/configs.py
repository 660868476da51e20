"""Workload shapes (plain data).

Shapes follow the paper's model settings (Table 1: N_res/N_seq/N_extra_seq =
256/128/1024 for initial training, 384/512 for fine-tuning) and the caption of
Table 5 (head=8, N_seq=128, N_res=256, C_m=256, C_z=128).  Head sizes, hidden
sizes and the transition factor are the AlphaFold2 values the paper defers to.
"""

_F32, _BF16 = 0, 1


def _dims(s, r, c_m, c_z, h_msa, d_msa, h_pair, d_pair, c_tri, c_opm,
          n_trans=4, col_global=0, dtype=_BF16, variant=0):
    # variant: 0 Parallel Evoformer (Figure 1(c)), 1 AlphaFold2 (1(a)), 2 AlphaFold-Multimer (1(b))
    return dict(s=s, r=r, c_m=c_m, c_z=c_z, h_msa=h_msa, d_msa=d_msa,
                h_pair=h_pair, d_pair=d_pair, c_tri=c_tri, c_opm=c_opm,
                n_trans=n_trans, col_global=col_global, dtype=dtype,
                ln_eps=1e-5, opm_eps=1e-3, variant=variant)


# name -> (dims, mask recipe, seed)
CONFIGS = {
    # tiny fp32 block: last 3 residues masked
    "tiny": (_dims(8, 16, 32, 16, 4, 8, 2, 8, 16, 8, dtype=_F32),
             ("last_residues", 3), 0),
    # AF2 initial-training block
    "af2_initial": (_dims(128, 256, 256, 128, 8, 32, 4, 32, 128, 32),
                    ("random_residues", 0.10), 1),
    # extra-MSA-stack block (global column attention)
    "extra_msa": (_dims(1024, 256, 64, 128, 8, 8, 4, 32, 128, 32, col_global=1),
                  ("random_rows", 0.05), 2),
    # AF2 fine-tuning-shape block
    "af2_finetune": (_dims(512, 384, 256, 128, 8, 32, 4, 32, 128, 32),
                     ("random_residues", 0.10), 3),
    # extra-MSA-stack block at the fine-tuning depth (Table 1: N_extra_seq 5120, N_res 384);
    # too large for the float64 oracle: timed, and tested through size-independent properties
    "extra_msa_finetune": (_dims(5120, 384, 64, 128, 8, 8, 4, 32, 128, 32, col_global=1),
                           ("random_rows", 0.05), 6),
}

# a very small shape for brute-force loops and finite differences
TINY_TEST_DIMS = _dims(3, 4, 8, 8, 2, 4, 2, 4, 4, 2, n_trans=2, dtype=_F32)


def dims_for(name):
    d, mask, seed = CONFIGS[name]
    return dict(d), mask, seed
