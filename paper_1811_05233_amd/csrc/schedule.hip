// Host-side training-recipe functions of the paper's configuration B and its batch-size control table
// (Sec. 3.2 "Training Configurations", the three printed formulas, and Table 3).  Pure functions: they feed
// rn50_hparams (lr, momentum) and the per-GPU batch of rn50_config from one step to the next; nothing here
// touches the device.
#include "common.h"

// epoch = processed samples / data-set size (a real number in [0, 90])
extern "C" double rn50_sched_lr_b(double epoch)
{
    if (epoch < 5.0) return 0.2 + (29.0 - 0.2) * epoch / 5.0;          // 5-epoch warm-up
    const double d = 1.0 - epoch / 90.0;
    return (epoch < 30.0 ? 29.0 : 50.0) * d * d;                       // base LR 29, then 50, squared decay to epoch 90
}

extern "C" double rn50_sched_noise_scale_b(double epoch) { return rn50_sched_lr_b(epoch) * 32.0 * 1024.0 / (1.0 - 0.9); }

// total_batch = total mini-batch size over all GPUs.  Where the learning rate is zero (epoch 90) the ratio
// LR/NoiseScale is taken at its constant value (1 - 0.9)/(32*1024).
extern "C" double rn50_sched_momentum_b(double epoch, double total_batch)
{
    const double lr = rn50_sched_lr_b(epoch);
    if (lr == 0.0) return 1.0 - total_batch * (1.0 - 0.9) / (32.0 * 1024.0);
    return 1.0 - lr * total_batch / rn50_sched_noise_scale_b(epoch);
}

// Table 3: per-worker and total mini-batch size of experiment `experiment` (0 = Reference, 1..4 = Exp. 1..4) at
// `epoch` (columns: the first 30 epochs, up to 45, up to 75, up to 90; "K" = 1024).  RN50_ERR_SHAPE for an
// unknown experiment or an epoch outside [0, 90].
extern "C" int rn50_sched_batch(int experiment, double epoch, int* per_worker, int* total)
{
    if (!per_worker || !total) return RN50_ERR_NULL;
    if (experiment < 0 || experiment > 4 || !(epoch >= 0.0) || epoch > 90.0) return RN50_ERR_SHAPE;
    const int col = epoch < 30.0 ? 0 : epoch < 45.0 ? 1 : epoch < 75.0 ? 2 : 3;
    static const int worker[5][4] = {{32, 32, 32, 32}, {16, 32, 32, 32}, {16, 32, 32, 32}, {16, 32, 32, 32}, {16, 16, 32, 32}};
    static const int total_k[5][4] = {{32, 32, 32, 32}, {34, 68, 68, 68}, {54, 54, 54, 54}, {54, 64, 64, 64}, {34, 68, 85, 119}};
    *per_worker = worker[experiment][col];
    *total = total_k[experiment][col] * 1024;
    return RN50_OK;
}
