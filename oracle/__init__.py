"""CPU checker for the multiplexed-module hot path.  Test infrastructure only: the
product package never imports it."""
