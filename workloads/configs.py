"""The five benchmark configurations: teacher and student shapes, batch sizes, unroll."""
from .nets import mlp, nature_cnn, impala_cnn, paper_small_cnn

CONFIGS = {
    # classic-control MLP: same shape for teacher (fp32) and student (int8)
    0: dict(name="classic_mlp", teacher=mlp("classic_mlp_t", 4, (64, 64), 2),
            student=mlp("classic_mlp_s", 4, (64, 64), 2), teacher_precision="fp32",
            student_from="quantize", batches=(32,), calib=256),
    # Box2D-style MLP: wide fp32 teacher, independently initialised narrow int8 student
    1: dict(name="box2d_mlp", teacher=mlp("box2d_mlp_t", 24, (256, 256), 4),
            student=mlp("box2d_mlp_s", 24, (64, 64), 4), teacher_precision="fp32",
            student_from="independent", batches=(1024, 8192), calib=256),
    # Nature-DQN CNN on Atari-like frames: bf16 teacher, int8 student of the same shape
    2: dict(name="nature_cnn", teacher=nature_cnn("nature_cnn_t"), student=nature_cnn("nature_cnn_s"),
            teacher_precision="bf16", student_from="quantize", batches=(160, 4096), calib=256),
    # IMPALA deep ResNet: bf16 teacher, 50 % channel-pruned int8 student
    3: dict(name="impala_resnet", teacher=impala_cnn("impala_t", (16, 32, 32)),
            student=impala_cnn("impala_s", (8, 16, 16)), teacher_precision="bf16",
            student_from="prune", batches=(160, 1024, 16384), calib=256),
    # IMPALA CNN + LSTM core, unrolled 16 steps
    4: dict(name="impala_lstm", teacher=impala_cnn("impala_lstm_t", (16, 32, 32), lstm_hidden=256),
            student=impala_cnn("impala_lstm_s", (8, 16, 16), lstm_hidden=256), teacher_precision="bf16",
            student_from="prune", batches=(4096,), calib=256, unroll=16),
}

# the compressed networks of the paper's own network table (two convs, small FC)
PAPER_STUDENTS = {
    "net1": paper_small_cnn("net1", 16, 32, 256),
    "net2": paper_small_cnn("net2", 8, 16, 128),
    "net3": paper_small_cnn("net3", 4, 4, 32),
}


def get_config(i):
    return CONFIGS[int(i)]
