"""Learning-rate schedule of the paper's BERT-Large seqlen-128 run (Section 6, "Training
parameters"), used as a per-step input by the two-stage driver tests: the rate starts at lr0, grows
exponentially to lr_peak over the first `rampup` steps, then is multiplied by `decay` after every
`decay_every` further steps.  The paper's values: lr0 = 1e-3, lr_peak = 12e-3, rampup = 450,
decay = 0.9 every 250 steps, 5993 steps in all, the first 1000 (16.7 %) being the LAMB warmup stage.
"""


def lr_seqlen128(t, lr0=1e-3, lr_peak=12e-3, rampup=450, decay=0.9, decay_every=250):
    if t < rampup:
        return lr0 * (lr_peak / lr0) ** (t / float(rampup))
    return lr_peak * decay ** ((t - rampup) // decay_every)


PAPER_SEQLEN128 = dict(total_steps=5993, warmup_steps=1000)
PAPER_SEQLEN512 = dict(total_steps=555, warmup_steps=107)
