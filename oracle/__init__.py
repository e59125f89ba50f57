"""CPU oracle of the AutoAssist shrink + SGD path.  TEST INFRASTRUCTURE ONLY."""
