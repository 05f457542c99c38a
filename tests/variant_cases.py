"""Problem sizes (classes C, padded target length Lmax) that between them make w2l_ctc_fwd_bwd and
w2l_asg_fwd_bwd launch every variant of their lattice kernels; which variant a size takes is asked
of the library's own host-side query (w2l_ctc_launch_config / w2l_asg_launch_config), the function
the entry points dispatch through."""

# CTC: (pairs per lane, frames per block) follows Lmax + 1 pairs: <= 208 -> (1,16), <= 220 -> (1,12),
# <= 416 -> (2,16), <= 440 -> (2,12), <= 832 -> (4,16), <= 880 -> (4,12), more -> (4,16) on more wavefronts;
# the score-table values per thread follow frames per block * C against the workgroup size.
CTC_LMAX = [200, 215, 400, 436, 800, 870, 1100]
CTC_CLASSES = [29, 50, 100, 200]
CTC_CASES = [(c, l) for l in CTC_LMAX for c in CTC_CLASSES] + [(29, 60), (600, 20)]

# ASG: positions per lane / frames per block follow Lmax the same way (without the +1); 32 or 64 class
# lanes follow C; emission values staged per thread follow frames per block * C against the workgroup size.
ASG_CASES = [(c, l) for l in [90, 190, 205, 300, 380, 412, 500, 760, 828, 1100] for c in [8, 28, 40, 64]] + [(28, 250)]


def ctc_variant(P, C, Lmax):
    ppt, nq, blk, _ = P.w2l_ctc_launch_config(C, Lmax)
    return (ppt, nq, blk)


def asg_variant(P, C, Lmax):
    ppt, cmax, maxt, blk, nq, _ = P.w2l_asg_launch_config(C, Lmax)
    return (ppt, cmax, maxt, blk, nq)
