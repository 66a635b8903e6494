"""Training recipe of the paper's configuration B and Table 3 -- TEST INFRASTRUCTURE ONLY.

Plain definitions written from Sec. 3.2 ("Training Configurations": the three printed formulas for the
learning rate, the noise scale and the momentum) and from Table 3 (mini-batch size per worker and in total,
per range of epochs; "K" = 1024).  epoch = processed samples / data-set size."""


def lr_b(epoch):
    if epoch < 5:
        return 0.2 + (29 - 0.2) * epoch / 5
    if epoch < 30:
        return 29 * (1 - epoch / 90) ** 2
    return 50 * (1 - epoch / 90) ** 2


def noise_scale_b(epoch):
    return lr_b(epoch) * 32 * 1024 / (1 - 0.9)


def momentum_b(epoch, total_batch):
    return 1 - lr_b(epoch) * total_batch / noise_scale_b(epoch)


# experiment -> [(first epoch of the range, per worker, total in K)], ranges as the table's columns
TABLE3 = {
    0: [(0, 32, 32)],
    1: [(0, 16, 34), (30, 32, 68)],
    2: [(0, 16, 54), (30, 32, 54)],
    3: [(0, 16, 54), (30, 32, 64)],
    4: [(0, 16, 34), (30, 16, 68), (45, 32, 85), (75, 32, 119)],
}


def batch(experiment, epoch):
    row = [r for r in TABLE3[experiment] if epoch >= r[0]][-1]
    return row[1], row[2] * 1024
