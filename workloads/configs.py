"""The five benchmark configurations (synthetic stand-ins shaped like the paper's workloads).

Config 2 is shaped like the binary density-estimation sets / binarised 28x28
digits of Sec. 4.1, config 3 like 28x28 grey images, config 4 like the 32x32x3
street-number images and config 5 like a 64x64x3 crop of the face images of
Sec. 4.2.  None of those datasets is used: every sample is drawn from a seeded
mixture, see generate.py.
"""
BERNOULLI = 0
GAUSSIAN = 1
BINOMIAL = 2
CATEGORICAL = 3

CONFIGS = [
    dict(
        name="cfg1_rat_d8_k4",
        structure=dict(kind="rat", D=8, depth=3, R=2),
        K=4, channels=1, family=BERNOULLI, B=64,
        leaf_range=(0.1, 0.9),
        data=dict(kind="bernoulli_iid", p=0.5),
        mask=None,
    ),
    dict(
        name="cfg2_rat_d784_k10",
        structure=dict(kind="rat", D=784, depth=8, R=10),
        K=10, channels=1, family=BERNOULLI, B=100,
        leaf_range=(0.05, 0.95),
        data=dict(kind="bernoulli_mixture", components=10, lo=0.05, hi=0.95),
        mask=None,
    ),
    dict(
        name="cfg3_pd_28x28_k16",
        structure=dict(kind="pd", H=28, W=28, deltas=[7], axes=3),
        K=16, channels=1, family=GAUSSIAN, B=256,
        leaf_range=(0.0, 1.0),
        data=dict(kind="gaussian_mixture", components=20, std=0.1),
        mask=dict(kind="shared", observed_fraction=0.7),
    ),
    dict(
        name="cfg4_pd_32x32x3_k40",
        structure=dict(kind="pd", H=32, W=32, deltas=[8], axes=3),
        K=40, channels=3, family=GAUSSIAN, B=128,
        leaf_range=(0.0, 1.0),
        data=dict(kind="gaussian_mixture", components=50, std=0.1),
        mask=None,
    ),
    dict(
        name="cfg5_pd_64x64x3_k20",
        structure=dict(kind="pd", H=64, W=64, deltas=[16, 8], axes=3),
        K=20, channels=3, family=GAUSSIAN, B=64,
        leaf_range=(0.0, 1.0),
        data=dict(kind="gaussian_mixture", components=100, std=0.1),
        mask=dict(kind="shared", observed_fraction=0.5),
    ),
]


def get_config(i):
    """i is 1-based, as in the configuration list."""
    return CONFIGS[i - 1]


def fig3_config(K=10, depth=4, R=10, B=100):
    """One point of the efficiency sweeps of Sec. 4.1 (Fig. 3 and the inference-time figure of App. C):
    random binary trees over D = 512 variables of Gaussian noise, one-dimensional Gaussian leaves,
    defaults depth 4, R 10, K 10; inference is timed on batches of 100."""
    return dict(
        name=f"fig3_rat_d512_depth{depth}_r{R}_k{K}",
        structure=dict(kind="rat", D=512, depth=depth, R=R),
        K=K, channels=1, family=GAUSSIAN, B=B,
        leaf_range=(-1.0, 1.0),
        data=dict(kind="gaussian_noise"),
        mask=None,
    )


def sec42_config(shape="svhn"):
    """One mixture component of the image experiments of Sec. 4.2: Poon-Domingos structure with vertical
    splits only, four strips (step 8 on 32x32, step 32 on 128x128), K = 40, Gaussian leaves factorised
    over the three colour channels, mini-batches of 500.  Stand-in data: a seeded Gaussian mixture in
    [0, 1], not the street-number or face images."""
    H, delta = {"svhn": (32, 8), "celeba": (128, 32)}[shape]
    return dict(
        name=f"sec42_{shape}_pd_{H}x{H}x3_k40",
        structure=dict(kind="pd", H=H, W=H, deltas=[delta], axes=2),
        K=40, channels=3, family=GAUSSIAN, B=500,
        leaf_range=(0.0, 1.0),
        data=dict(kind="gaussian_mixture", components=5, std=0.1),
        mask=None,
        em=dict(step=0.5, min_var=1e-6, max_var=1e-2, w_floor=1e-9),
    )
